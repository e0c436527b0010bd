"""MI355X-native ranking hot path of arXiv 1407.4764 (on-the-fly category retrieval).

`paper_1407_4764_amd.binding` exposes the C-ABI entry points of libotf (hand-written HIP
for gfx950); `paper_1407_4764_amd.synth` draws the seeded synthetic inputs.  Importing the
package loads nothing; the shared library is opened on first use of the binding and a
missing library is an error, never a silent fallback.
"""
__all__ = ["binding", "synth"]
