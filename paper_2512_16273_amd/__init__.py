"""MI355X-native hot path of Truncated Sparse Logits Transmission (TSLT).

`paper_2512_16273_amd.tslt` is the thin binding over the C-ABI library built from `csrc/`;
`paper_2512_16273_amd.workloads` makes the seeded synthetic inputs.  Nothing is loaded at
package import: the HIP library is opened on first use and its absence is an error.
"""
