"""MI355X-native population step of Population Based Training.

`binding` wraps the C-ABI library built from `csrc/`; `workloads` names the
synthetic workloads and draws their seeded inputs.  Nothing is loaded at import
time; the library is opened on first use and its absence is an error.
"""
