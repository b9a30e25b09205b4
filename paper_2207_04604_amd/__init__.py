"""MI355X-native hot path of D2-MHE's private gradient exchange (multiparty BFV in RNS form).

``paper_2207_04604_amd.binding`` is the thin Python front-end of the C-ABI HIP library;
``paper_2207_04604_amd.synth`` holds the seeded synthetic workloads.
"""
