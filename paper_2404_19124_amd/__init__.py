"""MI355X-native draft + verify step of the combined token/embedding speculator
(arXiv 2404.19124).  The compute lives in the HIP library under csrc/ behind the
C ABI declared in include/spec.h; `binding` marshals arguments to it and
`workloads` draws seeded synthetic inputs.  Importing the package loads nothing
native; the binding raises if the built library is missing."""
__all__ = ["binding", "workloads"]
