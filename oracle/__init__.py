"""TEST INFRASTRUCTURE — the CPU oracle and the offline compressor the HIP library is checked
against.  Never imported by the product path."""
