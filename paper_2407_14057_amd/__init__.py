"""MI355X-native pruned prefill (LazyLLM, arxiv 2407.14057): C-ABI library + thin binding.

`binding` marshals arguments into liblazyllm.so; `synth` draws the seeded inputs;
`build` compiles the library.  Nothing is imported eagerly so that the input generators
can be used without the library being present.
"""
