"""MI355X-native MoE expert-layer library (gate, workload histogram, residual-based workload prediction,
masked grouped SwiGLU expert FFN, weighted combine) behind a C ABI; see include/moe_layer.h.

``paper_2602_03495_amd.workloads`` draws synthetic inputs (numpy only, importable without a GPU);
``paper_2602_03495_amd.binding`` marshals torch device tensors into the C ABI and needs the built library.
"""
