"""MI355X-native hot path of SAGE (entropy-guided adaptive speculative decoding).

`paper_2602_00523_amd.sage` binds the C-ABI HIP library (four calls, same names);
`paper_2602_00523_amd.workloads` draws the seeded synthetic inputs.  Importing the
package does not load the library; calling into it without a built library raises.
"""
