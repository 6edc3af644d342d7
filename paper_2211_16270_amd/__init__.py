"""MI355X-native transducer joint -> loss -> gradient path (arxiv 2211.16270, Algorithm 1).

`paper_2211_16270_amd.binding` is the thin ctypes layer over the C-ABI library built from
`csrc/`; `paper_2211_16270_amd.synth` draws the seeded synthetic batches.  Importing the
package loads nothing native; the first call into the binding does, and raises if the
library has not been built."""
