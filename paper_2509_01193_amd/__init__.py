"""MI355X-native multi-adapter LoRA linear layer (forward + backward) over packed batches.

``paper_2509_01193_amd.binding`` wraps the C-ABI library built from ``csrc/``;
``paper_2509_01193_amd.workloads`` holds the seeded synthetic inputs.  Importing the
package itself loads nothing native, so CPU-only tools can use the workloads.
"""
__all__ = ["binding", "workloads", "build"]
