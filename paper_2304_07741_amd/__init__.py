"""MI355X-native executor for Canvas micro-DAG kernels (forward and backward).

`binding` wraps the C-ABI library (`canvas_dag_compile`, `canvas_dag_forward`,
`canvas_dag_backward`, ...); `workloads` generates the seeded synthetic inputs.
Importing the package does not load the HIP library; the first call through
`binding` does, and raises if it has not been built.
"""
