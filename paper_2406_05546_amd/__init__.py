"""MI355X-native parameter-server hot path of arxiv 2406.05546 (worker CNN gradients on stale
snapshots + sync / async / stateless-buffered apply).  The HIP library is loaded on first use of
`binding`; importing the package itself (e.g. for `synth`) does not need it."""

__all__ = ["binding", "synth", "replay"]
