"""dbsn: on-line back-propagation for big plain MLPs and on-the-fly image
deformation, hand-written for MI355X (gfx950).

`paper_1003_0358_amd.binding` wraps the C-ABI library (include/dbsn.h);
`paper_1003_0358_amd.datagen` makes the seeded synthetic inputs.  Importing the
package loads nothing; `binding.load()` raises if the HIP library is not built.
"""
