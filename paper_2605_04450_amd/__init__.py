"""MI355X-native hot path of an HSTU serving step over one shared EMB/KV page pool.

`paper_2605_04450_amd.binding` wraps the C-ABI library (libracer_hip.so);
`paper_2605_04450_amd.synth` draws seeded synthetic workloads.  Importing the
package loads nothing: the library is opened on first use and its absence is
an error, never a fallback.
"""
