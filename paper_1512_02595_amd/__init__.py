"""Batched CTC loss and gradient for MI355X (gfx950), behind a C-ABI library.

`paper_1512_02595_amd.ctc` is the ctypes binding to the HIP library;
`paper_1512_02595_amd.workloads` draws the synthetic batches.  Importing the
package does not load the library; the binding does so on first use and raises
if it has not been built.
"""
__all__ = ["ctc", "workloads"]
