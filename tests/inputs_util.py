"""Input preparation shared by the tests (no expected values come from here): float inputs made
from un-deformed uint8 images, handed to the library and to the oracle alike."""
import numpy as np


def pixels_to_inputs(images_u8):
    """uint8 intensities -> float32 inputs in [-1, 1]."""
    return (images_u8.astype(np.float32) / np.float32(127.5) - np.float32(1.0)).astype(np.float32)
