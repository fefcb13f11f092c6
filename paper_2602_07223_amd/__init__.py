"""MI355X-native verify -> select -> draft attention path of Vegas (verification-guided sparse attention).

``paper_2602_07223_amd.binding`` loads the HIP library and exposes the three C-ABI calls;
``paper_2602_07223_amd.synth`` draws the seeded synthetic workloads.  Importing this package does not
load the library: that happens on first use of the binding and fails loudly if it is not built.
"""
__all__ = ["binding", "synth", "build"]
