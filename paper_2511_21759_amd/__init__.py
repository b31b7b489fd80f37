"""MI355X-native block-decode step and cache-refresh prefill of ODB-dLLM.

`paper_2511_21759_amd.binding` wraps the C-ABI library (include/odb.h);
`paper_2511_21759_amd.workloads` draws the seeded synthetic inputs.  Importing
this package loads neither: the HIP library is opened on first use and its
absence is an error, never a fallback.
"""
