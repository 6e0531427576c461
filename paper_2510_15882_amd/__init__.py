"""MI355X-native local share of FlexLink's AllReduce / AllGather.

The product is the C-ABI library built from csrc/ (see include/flexlink.h);
`binding` marshals torch tensors into it and `workloads` generates the seeded
synthetic inputs.  Nothing is imported eagerly so that `workloads` can be used
without the built library.
"""
__all__ = ["binding", "workloads", "build"]
